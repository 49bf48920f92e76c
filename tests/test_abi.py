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
    # the static-workspace variant refuses what its 64 MiB array cannot hold, before anything else happens
    assert lib.ql_w8a8_linear_static(vp(0x1000), 11008, 16384, 11008, vp(0x2000), vp(0x3000), None, 4096, vp(0x4000),
                                     4096, None) == 5
    # unknown kernel variant
    assert lib.ql_set_kernel_variant(77) == 4
    assert lib.ql_set_kernel_variant(0) == 0


def test_header_is_plain_c_and_a_c_program_links(tmp_path):
    """The boundary is a C ABI: the header compiles as strict C99 and a C program that calls the host-only
    entry points links against the library and runs (no GPU needed for these calls)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    lib_path = os.path.join(ROOT, "paper_2512_23367_amd", "libqlinear.so")
    if not os.path.exists(lib_path):
        pytest.skip("library not built")
    src = tmp_path / "use_abi.c"
    src.write_text(
        '#include <stdio.h>\n#include "qlinear.h"\n'
        "int main(void) {\n"
        "    size_t canon = 0, scales = 0, kernel = 0, ws = 0;\n"
        "    int block = 0;\n"
        "    ql_plan plan;\n"
        "    if (ql_version() < 100) return 1;\n"
        "    if (ql_weight_bytes(4096, 4096, 4, 128, &canon, &scales, &kernel) != QL_OK) return 2;\n"
        "    if (canon != (size_t)4096 * 2048 || scales != (size_t)4096 * 32 * 2 || kernel < canon + 2 * scales) return 3;\n"
        "    if (ql_workspace_bytes(64, 512, 512, 8, &ws) != QL_OK || ws < (size_t)64 * 512) return 4;\n"
        "    if (ql_hadamard_block(11008, &block) != QL_OK || block != 256) return 5;\n"
        "    if (ql_weight_bytes(10, 100, 8, 0, &canon, &scales, &kernel) != QL_ERR_SHAPE) return 6;\n"
        '    if (ql_last_error()[0] == 0) return 7;\n'
        "    if (ql_plan_gemm(1, 4096, 4096, 8, 0, 0, &plan) != QL_OK || plan.family != QL_FAMILY_DECODE) return 8;\n"
        "    if (ql_plan_gemm(4096, 4096, 4096, 8, 0, 0, &plan) != QL_OK || plan.family != QL_FAMILY_TILE || plan.est_us <= 0) return 9;\n"
        '    printf("ok %d\\n", ql_version());\n'
        "    return 0;\n}\n")
    exe = tmp_path / "use_abi"
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe), lib_path,
                    "-Wl,-rpath," + os.path.dirname(lib_path)], check=True, capture_output=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0 and out.stdout.startswith("ok"), (out.returncode, out.stdout, out.stderr)
