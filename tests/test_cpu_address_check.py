"""Address check of the HIP kernels without a GPU.

The library's sources are compiled for the host against a stand-in for the HIP runtime (tests/cpu_build/) and every
entry point is run thread by thread under AddressSanitizer and the alignment sanitizer on buffers that end where their
allocation ends: the real
index arithmetic of every kernel and of the host-side launch code is executed, and any access outside a buffer is
reported.  (Matrix-core products and LDS contents are stubs: results are not checked here, only addresses.)
The shapes include the full-size workloads of bench.py's extra legs and stacked / ragged backward passes at sizes the
GPU parity tests do not reach.
"""
import os
import re
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
CSRC = ROOT / "paper_2503_12211_amd" / "csrc"
CLANG = Path(os.environ.get("STL_HOST_CLANG", "/opt/rocm/llvm/bin/clang++"))

pytestmark = pytest.mark.skipif(not CLANG.exists(), reason=f"{CLANG} not found")

DMA = ('asm volatile("s_mov_b32 m0, %1\\n\\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(l) : "memory", "m0");')


def _host_source(text: str) -> str:
    """The few GPU-only constructs of a kernel file in host form: dynamic LDS becomes a heap block of exactly the size the launch asked for, the LDS-DMA load a
    16-byte read the sanitizer can see whose LDS destination is checked against the dynamic LDS size of the launch, hardware
    waits and barriers nothing."""
    text = text.replace("extern __shared__ __align__(16) char smem[];", "char *smem = cpu_dyn_lds_ptr();")
    assert "global_load_lds_dwordx4 %0" not in text or DMA in text, "LDS-DMA statement changed: update the host form"
    text = text.replace(DMA, "cpu_touch16(g, l);")
    # LDS addresses count from the start of the dynamic array in the host form
    for macro in ("STL_LDS", "STL_LDS_PTR"):
        text = text.replace(f"(uint32_t)(uintptr_t){macro}(smem)", "0u")
    text = re.sub(r'asm volatile\("s_barrier" ::: "memory"\);', ";", text)
    text = re.sub(r'asm volatile\("s_waitcnt [^;]*;', ";", text)
    text = re.sub(r'asm volatile\("" : "\+v"\(\w+\)\);', ";", text)      # opaque-value fences
    text = text.replace('asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");',
                        "*reinterpret_cast<u32x4_t *>(p) = v;")               # write-through store: a plain store on the host
    left = [ln for ln in text.splitlines() if "asm volatile" in ln and 'asm volatile("" :::' not in ln]
    assert not left, f"unhandled inline assembly: {left}"
    if "STL_PIPELINE_STATIC_TICKETS" in text:
        text = "#define STL_PIPELINE_STATIC_TICKETS 1\n" + text
    return text.replace('#include "../../include/stl.h"', '#include "stl.h"')


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    work = tmp_path_factory.mktemp("cpu_build")
    for f in list(CSRC.glob("*.hip")) + list(CSRC.glob("*.h")):
        (work / f.name.replace(".hip", ".cpp")).write_text(_host_source(f.read_text()))
    shutil.copy(ROOT / "include" / "stl.h", work / "stl.h")
    shutil.copy(ROOT / "tests" / "cpu_build" / "driver.cpp", work / "driver.cpp")
    flags = ["-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address,alignment", "-fno-sanitize-recover=alignment",
             "-fno-omit-frame-pointer", "-Wno-everything",
             f"-I{ROOT / 'tests' / 'cpu_build'}", f"-I{work}"]
    objs, procs = [], []
    for src in sorted(work.glob("*.cpp")):
        obj = src.with_suffix(".o")
        objs.append(obj)
        procs.append((src, subprocess.Popen([str(CLANG), *flags, "-c", str(src), "-o", str(obj)], stdout=subprocess.PIPE,
                                            stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, f"{src.name}:\n{out[-3000:]}"
    exe = work / "address_check"
    res = subprocess.run([str(CLANG), "-fsanitize=address,alignment", *map(str, objs), "-o", str(exe)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]

    def run(*cases, expect_ok=True):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")
        r = subprocess.run([str(exe), *cases], capture_output=True, text=True, env=env, timeout=900)
        text = r.stdout + r.stderr
        if expect_ok:
            assert r.returncode == 0 and "ERROR: AddressSanitizer" not in text and "runtime error" not in text, text[-4000:]
            assert text.count("  ok") == len(cases), text[-2000:]
        return r.returncode, text
    return run


def test_planted_overflow_is_reported(checker):
    """The check itself: an output buffer 32 bytes short must be reported, in the kernel that writes it."""
    rc, text = checker("plant", expect_ok=False)
    assert rc != 0 and "heap-buffer-overflow" in text and "decode_mfma_kernel" in text


def test_core_path_addresses(checker):
    checker("bwd:512:256:384:32", "bwd:1024:1024:1024:49", "bwd:260:36:44:7", "f32,bwd:64:32:48:17",
            "fwd:1024:512:512:32:2", "fwd:1024:512:512:16:3", "fwd:8192:4096:256:8:0", "fwd:2048:1024:1024:32:4",
            "fwd:2340:256:1024:17:4",
            "mlp:1024:256:1024:24", "mlp:64:40:36:9", "ewb:256:384:24", "ewb:64:36:8", "f32,ewb:96:160:17")


def test_tall_matrix_stays_within_grid_limits(checker):
    """More than a million tile rows through the any-shape kernels (fp32 storage; bf16 with a tile count that no
    matrix-core kernel takes): every launch extent must stay within the device limits, which the stand-in runtime
    checks for every launch, and every access in bounds."""
    checker("f32,bwd:4200000:8:8:2", "bwd:4200000:4:12:3")
    # the shapes of the GPU parity test on tall matrices (tests/test_gpu_backward.py)
    checker("bwd:560000:32:32:8", "f32,bwd:560004:8:8:2", "bwd:560004:24:8:5")


def test_two_activation_addresses(checker):
    checker("aa:3:256:128:256:32", "aa:2:1024:640:768:16", "aa:5:72:40:56:49", "aa:2:36:20:28:7", "f32,aa:3:64:32:48:17",
            "aa:8:1024:1024:1024:32")


def test_ragged_row_addresses(checker):
    checker("ragged:8:197:256:512:32", "ragged:3:198:64:96:24", "ragged:5:39:96:160:49", "ragged:4:21:40:36:7",
            "ragged:1:5:32:32:16", "f32,ragged:3:13:24:20:11", "ragged:4:64:64:64:32", "ragged:64:197:768:1024:32")


def test_full_size_extra_workloads(checker):
    """The attention-scores and attention-values shapes (32 stacked problems) and a stacked square batch, forward and
    backward."""
    checker("aa:32:1024:128:1024:32", "aa:32:1024:1024:128:32", "aa:8:2048:2048:2048:32")
