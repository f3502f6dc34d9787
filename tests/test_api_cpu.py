"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2407_13885_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "attnw.h")

OK, E_NULL, E_SHAPE, E_DTYPE, E_UNSUP, E_ALIGN, E_ALIAS, E_LAUNCH = 0, -1, -2, -3, -4, -5, -6, -7
F32, BF16 = 0, 1


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        binding.build()
    return binding.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(attnw_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    declared = _declared_functions()
    assert set(declared) == set(binding.EXPORTS)
    out = subprocess.run(["nm", "-D", "--defined-only", binding.library_path()], capture_output=True, text=True,
                         check=True).stdout
    exported = {line.split()[-1] for line in out.splitlines() if " T " in line}
    for name in declared:
        assert name in exported, name
        assert getattr(lib, name) is not None


def test_version_and_status_strings(lib):
    assert binding.attnw_version() >= 100
    seen = {binding.attnw_status_string(s) for s in range(0, -8, -1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert binding.attnw_status_string(-99) == "unknown status"


# fake, suitably aligned, non-overlapping "device" addresses: validation never dereferences them
QA, KA, PA = 0x10000000, 0x20000000, 0x40000000


def test_fused_validation_order(lib):
    f = lib.attnw_fused
    assert f(QA, KA, PA, 1, 1, 128, 64, 0.125, 7, None) == E_DTYPE
    assert f(None, None, None, 1, 1, 128, 64, 0.125, 7, None) == E_DTYPE          # dtype before null
    assert f(QA, KA, PA, -1, 1, 128, 64, 0.125, BF16, None) == E_SHAPE
    assert f(QA, KA, PA, 1, 1, -5, 64, 0.125, BF16, None) == E_SHAPE
    assert f(None, KA, PA, 1, 1, 128, 64, 0.125, BF16, None) == E_NULL
    assert f(QA, None, PA, 1, 1, 128, 64, 0.125, BF16, None) == E_NULL
    assert f(QA, KA, None, 1, 1, 128, 64, 0.125, BF16, None) == E_NULL
    assert f(QA, KA, PA, 1 << 40, 1 << 40, 128, 64, 0.125, BF16, None) == E_SHAPE  # B*H overflows
    assert f(QA, KA, PA, 1 << 20, 1 << 20, 1 << 20, 64, 0.125, BF16, None) == E_SHAPE
    for d in (0, 8, 24, 100, 272, 512):
        assert f(QA, KA, PA, 1, 1, 128, d, 0.125, BF16, None) == E_UNSUP, d
    for d in (0, 2, 6, 30, 260, 512):            # fp32 rows are whole 16-byte chunks: multiples of 4
        assert f(QA, KA, PA, 1, 1, 128, d, 0.125, F32, None) == E_UNSUP, d
    assert f(QA, KA, PA, 1, 1, (1 << 30) + 1, 64, 0.125, BF16, None) == E_UNSUP
    assert f(QA + 2, KA, PA, 1, 1, 128, 64, 0.125, BF16, None) == E_ALIGN
    assert f(QA, KA + 8, PA, 1, 1, 128, 64, 0.125, BF16, None) == E_ALIGN
    assert f(QA, KA, PA + 4, 1, 1, 128, 64, 0.125, F32, None) == E_ALIGN
    # P overlapping Q / K: Q is 128*64*2 = 16384 bytes long
    assert f(QA, KA, QA + 16384 - 16, 1, 1, 128, 64, 0.125, BF16, None) == E_ALIAS
    assert f(QA, KA, KA, 1, 1, 128, 64, 0.125, BF16, None) == E_ALIAS
    assert f(QA, PA + 128 * 128 * 2 - 16, PA, 1, 1, 128, 64, 0.125, BF16, None) == E_ALIAS


def test_empty_problems_are_ok_and_touch_nothing(lib):
    assert lib.attnw_fused(None, None, None, 0, 4, 128, 64, 0.125, BF16, None) == OK
    assert lib.attnw_fused(None, None, None, 2, 0, 128, 64, 0.125, F32, None) == OK
    assert lib.attnw_fused(None, None, None, 2, 2, 0, 64, 0.125, F32, None) == OK
    assert lib.attnw_gemm_scores(None, None, None, 2, 2, 0, 64, 0.125, F32, None) == OK
    assert lib.attnw_softmax(None, None, 0, 128, BF16, None) == OK
    assert lib.attnw_softmax(None, None, 128, 0, F32, None) == OK


def test_gemm_scores_shares_the_rules(lib):
    g = lib.attnw_gemm_scores
    assert g(QA, KA, PA, 1, 1, 128, 64, 0.125, 2, None) == E_DTYPE
    assert g(QA, KA, None, 1, 1, 128, 64, 0.125, F32, None) == E_NULL
    assert g(QA, KA, PA, 1, 1, 128, 22, 0.125, F32, None) == E_UNSUP
    assert g(QA, KA, QA, 1, 1, 128, 64, 0.125, F32, None) == E_ALIAS


def test_attention_validation(lib):
    a = lib.attnw_attention
    VA, OA = 0x30000000, 0x50000000
    assert a(QA, KA, VA, OA, 1, 1, 256, 64, 0.125, 9, None) == E_DTYPE
    assert a(QA, KA, VA, OA, 1, -1, 256, 64, 0.125, BF16, None) == E_SHAPE
    assert a(None, None, None, None, 0, 1, 256, 64, 0.125, BF16, None) == OK
    assert a(QA, KA, None, OA, 1, 1, 256, 64, 0.125, BF16, None) == E_NULL
    assert a(QA, KA, VA, None, 1, 1, 256, 64, 0.125, BF16, None) == E_NULL
    assert a(QA, KA, VA, OA, 1, 1, 256, 272, 0.125, BF16, None) == E_UNSUP      # bf16: d a multiple of 16 up to 256
    assert a(QA, KA, VA, OA, 1, 1, 256, 24, 0.125, BF16, None) == E_UNSUP
    assert a(QA, KA, VA, OA, 1, 1, 256, 22, 0.125, F32, None) == E_UNSUP        # fp32: d a multiple of 4 up to 256
    assert a(QA, KA, VA, OA, 1, 1, 256, 260, 0.125, F32, None) == E_UNSUP
    assert a(QA, KA, VA + 4, OA, 1, 1, 256, 64, 0.125, F32, None) == E_ALIGN
    assert a(QA, KA, VA, VA, 1, 1, 256, 12, 0.125, F32, None) == E_ALIAS
    assert a(QA, KA, VA + 2, OA, 1, 1, 256, 64, 0.125, BF16, None) == E_ALIGN
    assert a(QA, KA, VA, VA, 1, 1, 256, 64, 0.125, BF16, None) == E_ALIAS
    assert a(QA, KA, VA, QA + 256 * 64 * 2 - 16, 1, 1, 256, 64, 0.125, BF16, None) == E_ALIAS


def test_softmax_validation(lib):
    s = lib.attnw_softmax
    assert s(QA, PA, 4, 4, -1, None) == E_DTYPE
    assert s(QA, PA, -4, 4, BF16, None) == E_SHAPE
    assert s(QA, PA, 4, -4, BF16, None) == E_SHAPE
    assert s(None, PA, 4, 4, BF16, None) == E_NULL
    assert s(QA, None, 4, 4, BF16, None) == E_NULL
    assert s(QA, PA, 1 << 40, 1 << 40, BF16, None) == E_SHAPE
    assert s(QA, PA, (1 << 31), 8, BF16, None) == E_UNSUP
    assert s(QA + 1, PA, 4, 4, BF16, None) == E_ALIGN
    assert s(QA, PA + 8, 4, 4, F32, None) == E_ALIGN
    assert s(QA, QA + 16, 4, 8, F32, None) == E_ALIAS          # partial overlap
    # S == P exactly (in place) passes validation; it is exercised on the GPU


def test_softmax_cast_validation(lib):
    s = lib.attnw_softmax_cast
    assert s(QA, PA, 4, 8, 5, BF16, None) == E_DTYPE
    assert s(QA, PA, 4, 8, F32, -2, None) == E_DTYPE
    assert s(QA, PA, -4, 8, F32, BF16, None) == E_SHAPE
    assert s(None, None, 0, 8, F32, BF16, None) == OK
    assert s(None, PA, 4, 8, F32, BF16, None) == E_NULL
    assert s(QA, PA + 4, 4, 8, F32, BF16, None) == E_ALIGN
    assert s(QA, QA, 4, 8, F32, BF16, None) == E_ALIAS            # in place needs equal types
    assert s(QA, QA + 64, 4, 8, F32, BF16, None) == E_ALIAS       # bf16 output inside the fp32 input
    assert s(QA, QA + 128, 4, 8, F32, BF16, None) != E_ALIAS      # directly behind it: no overlap


def test_scale_validation(lib):
    s = lib.attnw_scale
    assert s(QA, PA, 16, 0.5, 7, None) == E_DTYPE
    assert s(QA, PA, -1, 0.5, BF16, None) == E_SHAPE
    assert s(None, None, 0, 0.5, BF16, None) == OK
    assert s(None, PA, 16, 0.5, BF16, None) == E_NULL
    assert s(QA, None, 16, 0.5, F32, None) == E_NULL
    assert s(QA, PA, 1 << 62, 0.5, F32, None) == E_SHAPE
    assert s(QA + 2, PA, 16, 0.5, BF16, None) == E_ALIGN
    assert s(QA, QA + 16, 16, 0.5, BF16, None) == E_ALIAS       # partial overlap
    # X == Y exactly (in place) passes validation; it is exercised on the GPU


def test_binding_raises_with_status(lib):
    with pytest.raises(binding.AttnwError) as ei:
        binding.attnw_softmax(QA + 1, PA, 4, 4, BF16)
    assert ei.value.status == E_ALIGN and "aligned" in str(ei.value)


def test_header_is_plain_c_and_a_c_program_links(lib, tmp_path):
    """include/attnw.h compiled as C99 with warnings as errors; a C caller links against libattnw.so and gets
    the validation answers without any GPU (validation runs before the first HIP call)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler on this host")
    src = tmp_path / "caller.c"
    src.write_text(
        '#include "attnw.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "  int bad = attnw_softmax((void *)16, (void *)32, -1, 4, ATTNW_BF16, 0);\n"
        "  int empty = attnw_fused(0, 0, 0, 0, 1, 128, 64, 0.125f, ATTNW_F32, 0);\n"
        '  printf("%d %d %d %s\\n", bad, empty, attnw_version(), attnw_status_string(bad));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "caller"
    libdir = os.path.dirname(binding.library_path())
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-l:libattnw.so", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 3)
    assert int(out[0]) == E_SHAPE and int(out[1]) == OK and int(out[2]) >= 100 and "shape" in out[3]


def test_product_package_does_not_import_the_oracle():
    """The oracle is test infrastructure: nothing under the product package may use it."""
    pkg = os.path.join(ROOT, "paper_2407_13885_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".hpp", ".cpp", ".c")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), fn
                assert "attnw_oracle" not in text, fn
