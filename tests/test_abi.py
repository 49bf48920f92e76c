"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
argument validation returns the documented status codes (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

from paper_2512_23367_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    hdr = open(os.path.join(ROOT, "include", "qlinear.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return sorted(set(re.findall(r"\b(ql_[a-z0-9_]+)\s*\(", hdr)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 15
    lib = binding.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in qlinear.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_version_and_sizes():
    assert binding.ql_version() >= 100
    canon, scales, kern = binding.ql_weight_bytes(100, 256, 8, 0)
    assert (canon, scales, kern) == (100 * 256, 400, 128 * 256)
    canon, scales, kern = binding.ql_weight_bytes(100, 256, 4, 128)
    assert canon == 100 * 128 and scales == 100 * 2 * 2
    assert kern == 128 * 128 + 2 * 512               # padded codes + two 256-aligned copies of the fp16 group scales
    assert binding.ql_act_kernel_bytes(33, 128) == 64 * 128
    assert binding.ql_workspace_bytes(33, 100, 128, 8) >= 64 * 128 + 33 * 4


@pytest.mark.parametrize("args,status", [
    ((100, 100, 8, 0), 2),          # K not a multiple of 64
    ((100, 192, 4, 128), 2),        # K not a multiple of 128 for int4
    ((100, 256, 8, 128), 4),        # unsupported (bits, group)
    ((100, 256, 4, 64), 4),
    ((0, 256, 8, 0), 2),
    ((100, 262144, 8, 0), 4),       # K beyond the int32-safe limit
])
def test_shape_validation(args, status):
    with pytest.raises(binding.QlError) as e:
        binding.ql_weight_bytes(*args)
    assert e.value.status == status
    assert binding.ql_last_error() != ""


def test_null_and_alignment_validation_without_launch():
    lib = binding.lib()
    vp = ctypes.c_void_p
    # NULL x
    assert lib.ql_quant_act_per_token(None, 128, 4, 128, vp(256), None, vp(256), None) == 1
    # misaligned x, bad ldx
    assert lib.ql_quant_act_per_token(vp(0x1008), 128, 4, 128, vp(256), None, vp(256), None) == 3
    assert lib.ql_quant_act_per_token(vp(0x1000), 100, 4, 128, vp(256), None, vp(256), None) == 3
    # M == 0 is a no-op even with NULL buffers
    assert lib.ql_quant_act_per_token(None, 128, 0, 128, None, None, None, None) == 0
    assert lib.ql_w8a8_linear(None, 128, 0, 128, None, None, None, 64, None, 64, None, 0, None) == 0
    # workspace too small
    assert lib.ql_w8a8_linear(vp(0x1000), 128, 4, 128, vp(0x2000), vp(0x3000), None, 64, vp(0x4000), 64,
                              vp(0x5000), 16, None) == 5
    # ldy not a multiple of 8
    assert lib.ql_w8a8_gemm(vp(0x1000), vp(0x2000), 4, 128, vp(0x3000), vp(0x4000), None, 64, vp(0x5000), 68,
                            None, 0, None) == 3
    # unknown kernel variant
    assert lib.ql_set_kernel_variant(77) == 4
    assert lib.ql_set_kernel_variant(0) == 0
