"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2409_00822_amd as R

    if not os.path.exists(R.lib_path()):
        from paper_2409_00822_amd import build

        build.build()
    return R.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rtopk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rtopk_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"rtopk_rowwise", "rtopk_rowwise_exact", "rtopk_rowwise_u8", "rtopk_rowwise_exact_u8", "rtopk_rowwise_eps", "rtopk_rowwise_smallest", "rtopk_rowwise_exact_smallest",
            "rtopk_rowwise_f16", "rtopk_rowwise_exact_f16", "rtopk_rowwise_bf16", "rtopk_rowwise_exact_bf16", "rtopk_maxk_dense",
            "rtopk_status_string", "rtopk_version", "rtopk_max_m"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_version_limits_and_status_strings(lib):
    assert lib.rtopk_version() >= 100
    assert lib.rtopk_max_m() == 65536
    seen = set()
    for code in range(0, -8, -1):
        s = lib.rtopk_status_string(code)
        assert s and s != b"unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert lib.rtopk_status_string(-99) == b"unknown status"


def test_argument_errors_are_reported_before_any_launch(lib):
    p = 4096  # a non-null, aligned, never dereferenced "device pointer"
    f = lib.rtopk_rowwise
    fe = lib.rtopk_rowwise_exact
    assert f(p, 0, 256, 32, 8, p, p, None) == 0            # N == 0: nothing to do
    assert f(None, 0, 256, 32, 8, None, None, None) == 0   # ... even with null pointers
    assert f(None, 4, 256, 32, 8, p, p, None) == -1
    assert f(p, 4, 256, 32, 8, None, p, None) == -1
    assert f(p, 4, 256, 32, 8, p, None, None) == -1
    assert f(p, -1, 256, 32, 8, p, p, None) == -2
    assert f(p, 4, 0, 1, 8, p, p, None) == -2
    assert f(p, 4, 256, 0, 8, p, p, None) == -2
    assert f(p, 4, 256, 257, 8, p, p, None) == -2
    assert f(p, 4, 256, 32, -1, p, p, None) == -3
    assert f(p, 4, 65537, 32, 8, p, p, None) == -4
    assert fe(p, 4, 70000, 32, p, p, None) == -4
    assert f(p, 2 ** 31, 9000, 32, 8, p, p, None) == -2   # one workgroup per row beyond 8192 columns: 2^31 - 1 rows
    assert lib.rtopk_rowwise_smallest(p, 4, 65540, 32, 8, p, p, None) == -4
    assert lib.rtopk_rowwise_exact_smallest(p, 4, 65540, 32, p, p, None) == -4
    assert lib.rtopk_rowwise_u8(p, 4, 260, 32, 8, p, p, None) == -4
    assert lib.rtopk_rowwise_exact_u8(p, 4, 260, 32, p, p, None) == -4
    fz = lib.rtopk_rowwise_eps
    fz.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p,
                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert fz(p, 4, 256, 32, -1e-3, p, p, None, None) == -7
    assert fz(p, 4, 256, 32, float("nan"), p, p, None, None) == -7
    assert fz(p, 0, 256, 32, 0.5, None, None, None, None) == 0
    assert fz(p, 4, 256, 32, 0.5, p, p, p + 2, None) == -5
    assert fz(p, 4, 65540, 32, 0.5, p, p, None, None) == -4
    assert f(p + 2, 4, 256, 32, 8, p, p, None) == -5
    assert f(p, 4, 256, 32, 8, p + 1, p, None) == -5
    assert f(p, 4, 256, 32, 8, p, p + 2, None) == -5
    fd = lib.rtopk_maxk_dense
    assert fd(p, 0, 256, 32, -1, p, None) == 0
    assert fd(None, 4, 256, 32, -1, p, None) == -1
    assert fd(p, 4, 256, 32, 8, None, None) == -1
    assert fd(p, 4, 256, 300, 8, p, None) == -2
    assert fd(p, 4, 70000, 32, 8, p, None) == -4
    assert fd(p + 2, 4, 256, 32, 8, p, None) == -5
    assert fd(p, 4, 256, 32, 8, p + 3, None) == -5
    # rows stored in 16 bits: 2-byte alignment is enough for values, the other checks are shared
    for name in ("rtopk_rowwise_f16", "rtopk_rowwise_bf16"):
        h = getattr(lib, name)
        assert h(p + 2, 0, 256, 32, 8, p + 2, p, None) == 0
        assert h(None, 4, 256, 32, 8, p, p, None) == -1
        assert h(p + 1, 4, 256, 32, 8, p, p, None) == -5
        assert h(p, 4, 256, 32, 8, p + 1, p, None) == -5
        assert h(p, 4, 256, 32, -2, p, p, None) == -3
        assert h(p, 4, 256, 300, 8, p, p, None) == -2
        assert h(p, 4, 70000, 32, 8, p, p, None) == -4
    for name in ("rtopk_rowwise_exact_f16", "rtopk_rowwise_exact_bf16"):
        h = getattr(lib, name)
        assert h(p, 4, 70000, 32, p, p, None) == -4
        assert h(p, 4, 256, 0, p, p, None) == -2


def test_binding_refuses_host_tensors():
    import torch

    import paper_2409_00822_amd as R

    with pytest.raises(ValueError):
        R.rtopk_rowwise_exact(torch.zeros(4, 8), 2)


def test_generated_search_loops_are_current():
    # rtopk_search_loops.inc is committed so that a plain hipcc build needs no Python; it must be what
    # the generator writes today
    import importlib.util

    csrc = os.path.join(ROOT, "paper_2409_00822_amd", "csrc")
    spec = importlib.util.spec_from_file_location("gen_search_loops", os.path.join(csrc, "gen_search_loops.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    committed = open(os.path.join(csrc, "rtopk_search_loops.inc")).read()
    gen.main()  # rewrites the file only if it differs
    assert open(os.path.join(csrc, "rtopk_search_loops.inc")).read() == committed


def test_header_is_plain_c_and_links_from_c(tmp_path, lib):
    # the boundary is a C ABI: the header must compile as C99, and a C program must link against the
    # library and reach the host-only entry points
    import shutil
    import subprocess

    import paper_2409_00822_amd as R

    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_rtopk.c"
    src.write_text(
        '#include "rtopk.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "  if (rtopk_max_m() != 65536 || rtopk_version() < 100) return 1;\n"
        "  /* argument errors are reported on the host, before any launch */\n"
        "  if (rtopk_rowwise(0, 4, 256, 32, 8, 0, 0, 0) != RTOPK_ERR_NULL_POINTER) return 2;\n"
        "  if (rtopk_rowwise_exact((const float*)64, 4, 256, 300, (float*)64, (int32_t*)64, 0) != RTOPK_ERR_BAD_SHAPE) return 3;\n"
        "  if (rtopk_maxk_dense(0, 0, 256, 32, -1, 0, 0) != RTOPK_OK) return 4;\n"
        '  printf("%s\\n", rtopk_status_string(RTOPK_ERR_M_TOO_LARGE));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "use_rtopk"
    libdir = os.path.dirname(R.lib_path())
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                           "-o", str(exe), "-L", libdir, "-l:librtopk.so", "-Wl,-rpath," + libdir])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, (out.returncode, out.stderr)
    assert "row width" in out.stdout
