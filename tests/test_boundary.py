"""CPU-side checks of the C ABI: the library loads, exports what include/stl.h declares, and rejects
bad arguments before any launch (no GPU needed: validation happens on the host)."""
import re
from pathlib import Path

import pytest

import paper_2503_12211_amd as stl

ROOT = Path(__file__).resolve().parent.parent
FAKE = 0x1000  # a non-null "device pointer"; never dereferenced because validation fails first


def test_header_symbols_are_exported():
    header = (ROOT / "include" / "stl.h").read_text()
    declared = set(re.findall(r"\b(stl_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    exported = set(stl.exported_symbols())
    assert declared <= exported, declared - exported


def test_version_and_status_strings():
    assert "gfx950" in stl.stl_version()
    assert stl.stl_status_string(0) == "ok"
    assert stl.stl_status_string(3).startswith("workspace")


@pytest.mark.parametrize("kw,status", [
    (dict(m=254), 1), (dict(k=0), 1), (dict(n=-4), 1), (dict(r=0), 1), (dict(r=65), 1),
    (dict(t=8), 2), (dict(dtype=7), 2),
])
def test_invalid_problem_is_rejected(kw, status):
    base = dict(m=256, k=256, n=256, r=32, dtype=stl.STL_BF16, t=4)
    base.update(kw)
    prob = stl.Problem(**base)
    assert stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD) == 0
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 1 << 40, 0, stream=0)
    assert e.value.status == status
    with pytest.raises(stl.StlError):
        stl.stl_backward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, 0, FAKE, 1 << 40, stream=0)
    with pytest.raises(stl.StlError):
        stl.stl_encode_weight(prob, FAKE, FAKE, FAKE, stream=0)


def test_null_pointers_and_workspace():
    prob = stl.Problem(256, 256, 256, 32)
    need = stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD, stl.STL_FLAG_UNFUSED)
    assert need >= 2 * 32 * 64 * 64 * 2
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward(prob, None, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, need, stl.STL_FLAG_UNFUSED, stream=0)
    assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, need - 1, stl.STL_FLAG_UNFUSED, stream=0)
    assert e.value.status == 3 and "workspace" in str(e.value)
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, 0, stl.STL_FLAG_UNFUSED, stream=0)
    assert e.value.status == 3
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, need, 0x4000, stream=0)
    assert e.value.status == 2
    bneed = stl.stl_workspace_bytes(prob, stl.STL_OP_BACKWARD)
    with pytest.raises(stl.StlError) as e:
        stl.stl_backward(prob, FAKE, FAKE, FAKE, FAKE, None, None, None, FAKE, FAKE, FAKE, FAKE, 0, FAKE, bneed, stream=0)
    assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:
        stl.stl_backward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, 2, FAKE, bneed, stream=0)
    assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:
        stl.stl_backward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, FAKE, FAKE, 0, FAKE, bneed - 1, stream=0)
    assert e.value.status == 3


def test_workspace_grows_with_problem():
    a = stl.stl_workspace_bytes(stl.Problem(256, 256, 256, 32), stl.STL_OP_BACKWARD)
    b = stl.stl_workspace_bytes(stl.Problem(512, 256, 256, 32), stl.STL_OP_BACKWARD)
    assert 0 < a < b
    assert stl.stl_workspace_bytes(stl.Problem(256, 256, 256, 32), stl.STL_OP_ENCODE_WEIGHT) == 0


def test_block_resident_variants_reject_unsupported_shapes():
    for kw in (dict(r=49), dict(k=96), dict(n=40), dict(dtype=stl.STL_F32)):
        base = dict(m=256, k=256, n=256, r=32, dtype=stl.STL_BF16)
        base.update(kw)
        prob = stl.Problem(**base)
        for flag in (stl.STL_FLAG_EPILOGUE, stl.STL_FLAG_FUSED):
            with pytest.raises(stl.StlError) as e:
                stl.stl_forward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 1 << 40, flag, stream=0)
            assert e.value.status == 2
    prob = stl.Problem(256, 256, 256, 32)
    with pytest.raises(stl.StlError) as e:      # the fused variant never materialises Xhat
        stl.stl_forward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 1 << 40, stl.STL_FLAG_FUSED, stream=0)
    assert e.value.status == 2
    assert stl.stl_workspace_bytes(prob, stl.STL_OP_FORWARD, stl.STL_FLAG_FUSED) == 0


def test_pipelined_variant_rejects_what_the_header_excludes():
    """STL_FLAG_PIPELINED: bf16, r <= 32, k and n multiples of 256, n >= 1024, m >= 2048 -- anything else is refused before
    any launch (the pointers here are not device memory)."""
    ok = dict(m=2048, k=1024, n=1024, r=32, dtype=stl.STL_BF16)
    assert stl.stl_workspace_bytes(stl.Problem(**ok), stl.STL_OP_FORWARD, stl.STL_FLAG_PIPELINED) > 0
    for kw in (dict(r=33), dict(k=1024 + 128), dict(n=1024 + 64), dict(n=768), dict(m=2044), dict(m=1024), dict(dtype=stl.STL_F32)):
        prob = stl.Problem(**{**ok, **kw})
        with pytest.raises(stl.StlError) as e:
            stl.stl_forward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 1 << 40, stl.STL_FLAG_PIPELINED, stream=0)
        assert e.value.status == 2, kw


def test_layer_pair_argument_checks():
    """stl_mlp_forward / stl_recode: chaining, variant, pointer and workspace checks happen before any launch."""
    up = stl.Problem(512, 256, 1024, 24, stl.STL_BF16)
    down = stl.Problem(512, 1024, 256, 16, stl.STL_BF16)
    need = stl.stl_mlp_workspace_bytes(up, down, 0)
    planes = 2 * (24 * 128 * 64 + 24 * 128 * 256 + 16 * 128 * 256 + 16 * 128 * 64)
    assert need == planes
    # the two-launch form adds the hidden activation
    assert stl.stl_mlp_workspace_bytes(up, down, stl.STL_FLAG_UNFUSED) == planes + 2 * 512 * 1024
    # fp32 storage has no one-pass kernel: hidden buffer included
    up32, down32 = stl.Problem(512, 256, 1024, 24, stl.STL_F32), stl.Problem(512, 1024, 256, 16, stl.STL_F32)
    assert stl.stl_mlp_workspace_bytes(up32, down32, 0) == 2 * planes + 4 * 512 * 1024
    args = (FAKE,) * 8
    for bad_down in (stl.Problem(512, 512, 256, 16), stl.Problem(256, 1024, 256, 16), stl.Problem(512, 1024, 256, 16, stl.STL_F32)):
        assert stl.stl_mlp_workspace_bytes(up, bad_down, 0) == 0
        with pytest.raises(stl.StlError) as e:
            stl.stl_mlp_forward(up, bad_down, *args, FAKE, 1 << 40, 0, stream=0)
        assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:
        stl.stl_mlp_forward(up, down, *args, FAKE, need - 1, 0, stream=0)
    assert e.value.status == 3
    with pytest.raises(stl.StlError) as e:
        stl.stl_mlp_forward(up, down, *args, FAKE, 1 << 40, stl.STL_FLAG_FUSED, stream=0)
    assert e.value.status == 2
    with pytest.raises(stl.StlError) as e:
        stl.stl_mlp_forward(up, down, None, *args[1:], FAKE, 1 << 40, 0, stream=0)
    assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:          # two-launch recode without its scratch
        stl.stl_recode(up, down, FAKE, FAKE, FAKE, FAKE, None, stl.STL_FLAG_UNFUSED, stream=0)
    assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:
        stl.stl_recode(up32, down32, FAKE, FAKE, FAKE, FAKE, None, 0, stream=0)
    assert e.value.status == 1


def test_weight_encoding_backward_argument_checks():
    prob = stl.Problem(256, 256, 512, 32, stl.STL_BF16)
    need = stl.stl_workspace_bytes(prob, stl.STL_OP_ENCODE_WEIGHT_BACKWARD)
    assert need >= 2 * 32 * 64 * 128                       # holds a bf16 copy of the planes
    need32 = stl.stl_workspace_bytes(stl.Problem(256, 256, 512, 32, stl.STL_F32), stl.STL_OP_ENCODE_WEIGHT_BACKWARD)
    assert 0 < need32 < need                               # fp32 storage: partial sums only
    for args, status in (((None, FAKE, FAKE, FAKE, FAKE, 0, FAKE, 1 << 40), 1), ((FAKE, FAKE, None, FAKE, FAKE, 0, FAKE, 1 << 40), 1),
                         ((FAKE, FAKE, FAKE, FAKE, FAKE, 2, FAKE, 1 << 40), 1), ((FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, need - 1), 3),
                         ((FAKE, FAKE, FAKE, FAKE, FAKE, 0, None, 0), 3)):
        with pytest.raises(stl.StlError) as e:
            stl.stl_encode_weight_backward(prob, *args, stream=0)
        assert e.value.status == status


def test_misaligned_pointers_are_rejected():
    """Data pointers must be 16-byte aligned; the check comes before any launch."""
    prob = stl.Problem(256, 256, 256, 32, stl.STL_BF16)
    odd = FAKE + 8
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward(prob, odd, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 1 << 40, 0, stream=0)
    assert e.value.status == 1 and "aligned" in str(e.value)
    with pytest.raises(stl.StlError) as e:
        stl.stl_backward(prob, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, odd, FAKE, 0, FAKE, 1 << 40, stream=0)
    assert e.value.status == 1 and "aligned" in str(e.value)
    for fn, args in ((stl.stl_encode_weight, (FAKE, odd, FAKE)), (stl.stl_encode_activation, (FAKE, FAKE, odd)),
                     (stl.stl_plane_matmul, (odd, FAKE, FAKE))):
        with pytest.raises(stl.StlError) as e:
            fn(prob, *args, stream=0)
        assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:
        stl.stl_decode(prob, FAKE, FAKE, odd, 0, stream=0)
    assert e.value.status == 1


def test_plane_layout_helpers():
    """stl_plane_elems and the test-side converters agree with the layout the header states:
    element (p, I, J) at ((I / 64) * r + p) * 64 * Cc + (I % 64) * Cc + J."""
    import numpy as np
    import gpu_util
    assert stl.STL_PLANE_GROUP == 64
    assert stl.stl_plane_elems(100, 8, 3) == 3 * 128 * 8
    assert stl.stl_plane_elems(128, 5, 7) == 7 * 128 * 5
    r, R, Cc = 3, 100, 8
    a = np.arange(r * R * Cc, dtype=np.float64).reshape(r, R, Cc)
    flat = gpu_util.group_planes(a)
    assert flat.size == stl.stl_plane_elems(R, Cc, r)
    for (p, I, J) in [(0, 0, 0), (2, 63, 7), (1, 64, 0), (2, 99, 3)]:
        assert flat[((I // 64) * r + p) * 64 * Cc + (I % 64) * Cc + J] == a[p, I, J]
    assert np.array_equal(gpu_util.ungroup_planes(flat, r, R, Cc), a)


def test_two_activation_argument_checks():
    prob = stl.Problem(256, 64, 256, 32, stl.STL_BF16)
    F, B = stl.STL_OP_FORWARD, stl.STL_OP_BACKWARD
    fwd, bwd = stl.stl_aa_workspace_bytes(prob, 4, F), stl.stl_aa_workspace_bytes(prob, 4, B)
    # stacked planes of A, B and Yhat; the backward adds their three gradients
    planes_bytes = 2 * (stl.stl_plane_elems(4 * 64, 16, 32) + stl.stl_plane_elems(4 * 16, 64, 32) + stl.stl_plane_elems(4 * 64, 64, 32))
    assert planes_bytes < fwd < planes_bytes + 8192 and bwd > 2 * planes_bytes      # + two r x 16 slots for a transposed basis
    assert stl.stl_aa_workspace_bytes(prob, 8, F) > fwd
    assert stl.stl_aa_workspace_bytes(prob, 0, F) == 0 and stl.stl_aa_workspace_bytes(prob, 4, 7) == 0
    assert stl.stl_aa_workspace_bytes(prob, 1 << 20, F) == 0          # stacked rows beyond the cap
    ok = [FAKE] * 6 + [None] * 3
    for nb, args, ws, flags, status in ((0, ok, (FAKE, 1 << 40), 0, 1), (4, [None] + ok[1:], (FAKE, 1 << 40), 0, 1),
                                        (4, ok, (FAKE, fwd - 1), 0, 3), (4, ok, (None, 0), 0, 3),
                                        (4, ok, (FAKE, 1 << 40), 0x400, 2), (4, ok, (FAKE, 1 << 40), stl.STL_FLAG_FUSED, 2),
                                        (4, [FAKE + 4] + ok[1:], (FAKE, 1 << 40), 0, 1)):
        with pytest.raises(stl.StlError) as e:
            stl.stl_aa_forward(prob, nb, *args, *ws, flags, stream=0)
        assert e.value.status == status, (nb, args, ws, flags)
    okb = [FAKE] * 6 + [None] * 3 + [FAKE] * 5
    for nb, args, acc, ws, status in ((4, okb[:5] + [None] + okb[6:], 0, (FAKE, 1 << 40), 1), (4, okb, 2, (FAKE, 1 << 40), 1),
                                      (4, okb, 0, (FAKE, bwd - 1), 3), (-1, okb, 0, (FAKE, 1 << 40), 1)):
        with pytest.raises(stl.StlError) as e:
            stl.stl_aa_backward(prob, nb, *args, acc, *ws, stream=0)
        assert e.value.status == status
    with pytest.raises(stl.StlError) as e:                # the backward takes only the transposed-operand flag
        stl.stl_aa_backward(prob, 4, *okb, 0, FAKE, 1 << 40, stl.STL_FLAG_GELU, stream=0)
    assert e.value.status == 2


def test_ragged_argument_checks():
    """Images of 197 rows: m must be a multiple of the rows per image, the fold is required when rows % 4 != 0."""
    prob = stl.Problem(8 * 197, 256, 512, 32, stl.STL_BF16)
    F, B = stl.STL_OP_FORWARD, stl.STL_OP_BACKWARD
    fwd, bwd = stl.stl_ragged_workspace_bytes(prob, 197, F), stl.stl_ragged_workspace_bytes(prob, 197, B)
    planes_bytes = 2 * (stl.stl_plane_elems(8 * 50, 64, 32) + stl.stl_plane_elems(8 * 50, 128, 32))   # over the padded tile rows
    assert planes_bytes < fwd < planes_bytes + 8192 and bwd > 2 * planes_bytes
    assert stl.stl_ragged_workspace_bytes(prob, 196, F) == 0          # 8*197 is not a multiple of 196
    assert stl.stl_ragged_workspace_bytes(prob, 3, F) == 0
    assert stl.stl_ragged_workspace_bytes(prob, 197, 9) == 0
    ok = [FAKE] * 6 + [None, None]
    for rows, args, ws, status in ((196, ok, (FAKE, 1 << 40), 1), (3, ok, (FAKE, 1 << 40), 1),
                                   (197, ok[:4] + [None] + ok[5:], (FAKE, 1 << 40), 1),      # fold missing
                                   (197, ok[:5] + [None] + ok[6:], (FAKE, 1 << 40), 1),      # C missing
                                   (197, ok, (FAKE, fwd - 1), 3), (197, ok, (None, 0), 3),
                                   (197, ok[:4] + [FAKE + 4] + ok[5:], (FAKE, 1 << 40), 1)):
        with pytest.raises(stl.StlError) as e:
            stl.stl_ragged_forward(prob, rows, *args, *ws, stream=0)
        assert e.value.status == status, (rows, args, ws)
    okb = [FAKE] * 6 + [None, None] + [FAKE] * 5
    for rows, args, acc, ws, status in ((197, okb, 3, (FAKE, 1 << 40), 1), (197, okb, 0, (FAKE, bwd - 1), 3),
                                        (197, okb[:5] + [None] + okb[6:], 0, (FAKE, 1 << 40), 1), (200, okb, 0, (FAKE, 1 << 40), 1)):
        with pytest.raises(stl.StlError) as e:
            stl.stl_ragged_backward(prob, rows, *args, acc, *ws, stream=0)
        assert e.value.status == status
    # a divisible row count needs no fold: the same call passes validation up to the workspace check
    even = stl.Problem(8 * 196, 256, 512, 32, stl.STL_BF16)
    with pytest.raises(stl.StlError) as e:
        stl.stl_ragged_forward(even, 196, FAKE, FAKE, FAKE, FAKE, None, FAKE, None, None, None, 0, stream=0)
    assert e.value.status == 3


def test_forward_static_rejects_before_any_device_call():
    """stl_forward_static validates on the host: bad arguments, unknown flags and problems whose planes do not fit the
    built-in scratch are refused without touching a device."""
    small = stl.Problem(256, 256, 256, 32)
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward_static(small, None, FAKE, FAKE, FAKE, FAKE, 0, stream=0)
    assert e.value.status == 1
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward_static(small, FAKE, FAKE, FAKE, FAKE, FAKE + 4, 0, stream=0)
    assert e.value.status == 1 and "aligned" in str(e.value)
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward_static(small, FAKE, FAKE, FAKE, FAKE, FAKE, stl.STL_FLAG_FUSED, stream=0)
    assert e.value.status == 2
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward_static(stl.Problem(254, 256, 256, 32), FAKE, FAKE, FAKE, FAKE, FAKE, 0, stream=0)
    assert e.value.status == 1
    # largest that fits and smallest that does not: r * roundup(M, 64) * (K + N) * 2 bytes against 64 MiB
    fits = stl.Problem(4 * 1024, 2048, 2048, 32)
    assert stl.stl_workspace_bytes(fits, stl.STL_OP_FORWARD, stl.STL_FLAG_UNFUSED) == stl.STL_STATIC_SCRATCH_BYTES
    over = stl.Problem(4 * 1025, 2048, 2048, 32)
    assert stl.stl_workspace_bytes(over, stl.STL_OP_FORWARD, stl.STL_FLAG_UNFUSED) > stl.STL_STATIC_SCRATCH_BYTES
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward_static(over, FAKE, FAKE, FAKE, FAKE, FAKE, 0, stream=0)
    assert e.value.status == 3 and "built-in scratch" in str(e.value)
    header = (ROOT / "include" / "stl.h").read_text()
    assert "#define STL_STATIC_SCRATCH_BYTES ((size_t)64 << 20)" in header


def test_dimension_cap_is_the_documented_one():
    header = (ROOT / "include" / "stl.h").read_text()
    cap = int(re.search(r"#define STL_MAX_DIM (\d+)", header).group(1))
    assert cap == 65535 * 256
    assert stl.stl_workspace_bytes(stl.Problem(cap, 4, 4, 1), stl.STL_OP_FORWARD) > 0
    assert stl.stl_workspace_bytes(stl.Problem(cap + 4, 4, 4, 1), stl.STL_OP_FORWARD) == 0
    with pytest.raises(stl.StlError) as e:
        stl.stl_forward(stl.Problem(4, cap + 4, 4, 1), FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 1 << 40, 0, stream=0)
    assert e.value.status == 1
