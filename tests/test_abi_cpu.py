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
            "rtopk_maxk_backward", "rtopk_maxk_backward_u8", "rtopk_maxk_backward_gather", "rtopk_maxk_backward_gather_u8",
            "rtopk_status_string", "rtopk_version", "rtopk_max_m"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_version_limits_and_status_strings(lib):
    assert lib.rtopk_version() >= 100
    assert lib.rtopk_max_m() == 1 << 24
    seen = set()
    for code in range(0, -9, -1):
        s = lib.rtopk_status_string(code)
        assert s and s != b"unknown status"
        seen.add(s)
    assert len(seen) == 9
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
    assert f(p, 4, (1 << 24) + 1, 32, 8, p, p, None) == -4
    assert fe(p, 4, (1 << 24) + 4, 32, p, p, None) == -4
    assert f(p, 2 ** 31, 9000, 32, 8, p, p, None) == -2   # one workgroup per row beyond 8192 columns: 2^31 - 1 rows
    assert lib.rtopk_rowwise_smallest(p, 4, (1 << 24) + 4, 32, 8, p, p, None) == -4
    assert lib.rtopk_rowwise_exact_smallest(p, 4, (1 << 24) + 4, 32, p, p, None) == -4
    assert lib.rtopk_rowwise_u8(p, 4, 260, 32, 8, p, p, None) == -4
    assert lib.rtopk_rowwise_exact_u8(p, 4, 260, 32, p, p, None) == -4
    fz = lib.rtopk_rowwise_eps
    fz.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p,
                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert fz(p, 4, 256, 32, -1e-3, p, p, None, None) == -7
    assert fz(p, 4, 256, 32, float("nan"), p, p, None, None) == -7
    assert fz(p, 0, 256, 32, 0.5, None, None, None, None) == 0
    assert fz(p, 4, 256, 32, 0.5, p, p, p + 2, None) == -5
    assert fz(p, 4, (1 << 24) + 4, 32, 0.5, p, p, None, None) == -4
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


def test_overlapping_buffers_are_refused_on_the_host(lib):
    base = 1 << 20  # never dereferenced: the range check happens before any launch
    N, M, k = 4, 256, 32
    in_bytes, out_bytes = N * M * 4, N * k * 4
    f, fe = lib.rtopk_rowwise, lib.rtopk_rowwise_exact
    assert f(base, N, M, k, 8, base, base + (1 << 16), None) == -8                   # values on top of the input
    assert f(base, N, M, k, 8, base + in_bytes - 4, base + (1 << 16), None) == -8    # last input word shared
    assert fe(base, N, M, k, base + (1 << 16), base + (1 << 16) + out_bytes - 4, None) == -8  # the two outputs
    assert lib.rtopk_rowwise_u8(base, N, M, k, 8, base + (1 << 16), base + in_bytes - 1, None) == -8
    fz = lib.rtopk_rowwise_eps
    fz.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p,
                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert fz(base, N, M, k, 0.1, base + (1 << 16), base + (1 << 17), base + (1 << 16) + 8, None) == -8  # iteration output
    assert lib.rtopk_maxk_dense(base, N, M, k, -1, base + in_bytes - 16, None) == -8
    assert lib.rtopk_rowwise_f16(base, N, M, k, 8, base + N * M * 2 - 2, base + (1 << 16), None) == -8
    # adjacent buffers are fine as far as this check goes: the call proceeds to the launch, which a
    # machine without a GPU refuses (-6) and a machine with one accepts (0, on memory it must not touch --
    # so only try it where there is no GPU)
    import torch

    if not torch.cuda.is_available():
        assert f(base, N, M, k, 8, base + in_bytes, base + in_bytes + out_bytes, None) == -6
    # the backward edge
    b, g = lib.rtopk_maxk_backward, lib.rtopk_maxk_backward_gather
    far, far2 = base + (1 << 16), base + (1 << 17)
    assert b(far, far2, N, M, k, far + 8, None) == -8        # dense output over its own input
    assert b(far, far2, N, M, k, far2 - in_bytes + 4, None) == -8  # dense output over the columns
    assert g(base, far2, N, M, k, base + in_bytes - 4, None) == -8
    assert g(base, far, N, M, k, far + out_bytes - 4, None) == -8  # gathered values over the columns


def test_backward_argument_errors(lib):
    p, q, r = 1 << 20, 1 << 21, 1 << 22
    for name, u8 in (("rtopk_maxk_backward", False), ("rtopk_maxk_backward_u8", True),
                     ("rtopk_maxk_backward_gather", False), ("rtopk_maxk_backward_gather_u8", True)):
        f = getattr(lib, name)
        assert f(None, None, 0, 256, 32, None, None) == 0
        assert f(None, q, 4, 256, 32, r, None) == -1
        assert f(p, None, 4, 256, 32, r, None) == -1
        assert f(p, q, 4, 256, 32, None, None) == -1
        assert f(p, q, -1, 256, 32, r, None) == -2
        assert f(p, q, 4, 256, 0, r, None) == -2
        assert f(p, q, 4, 256, 257, r, None) == -2
        assert f(p, q, 4, 70000, 32, r, None) == -4
        assert f(p + 2, q, 4, 256, 32, r, None) == -5
        assert f(p, q, 4, 256, 32, r + 1, None) == -5
        if u8:
            assert f(p, q, 4, 300, 32, r, None) == -4
        else:
            assert f(p, q + 2, 4, 256, 32, r, None) == -5


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
        "  if (rtopk_max_m() != (1 << 24) || rtopk_version() < 100) return 1;\n"
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


def test_toolchain_is_the_one_the_inline_assembly_was_validated_with():
    # The kernels contain hand-written hazard padding (s_nop after cross-lane writes and after 128-bit
    # stores issued from asm blocks) and EXEC-masked store blocks whose correctness depends on how this
    # compiler schedules around volatile asm.  They were validated (GPU parity suite, incl. the dense
    # M = 8192 regression) with the hipcc below; a different compiler must re-run that suite before this
    # pin is moved.
    import shutil
    import subprocess

    if shutil.which("hipcc") is None:
        pytest.skip("no hipcc")
    out = subprocess.run(["hipcc", "--version"], capture_output=True, text=True).stdout
    validated = ("HIP version: 7.2.", "roc-7.2.0")
    assert all(v in out for v in validated), (
        "hipcc differs from the validated toolchain (HIP 7.2 / roc-7.2.0 clang): re-run `pytest -m gpu` on an "
        "MI355X, then update this pin.\n" + out)


def test_every_expected_kernel_family_is_in_the_built_library():
    # a guard against an instantiation table silently losing a family: the symbol table of the built
    # library must name each kernel template and the shapes the headline paths dispatch to
    import shutil
    import subprocess

    import paper_2409_00822_amd as R

    if shutil.which("nm") is None:
        pytest.skip("no nm")
    if not os.path.exists(R.lib_path()):
        pytest.skip("library not built")
    syms = subprocess.run(["nm", "-D", "--defined-only", "-C", R.lib_path()], capture_output=True, text=True).stdout
    for needle in ("rtopk::rtopk_wave_kernel<4, 1, 4, true, 1, false, int, 0>",      # headline, exact
                   "rtopk::rtopk_wave_kernel<4, 1, 4, true, 0, false, int, 0>",      # headline, early stop
                   "rtopk::rtopk_wave_kernel<4, 1, 2, true, 1, false, unsigned char, 0>",  # few rows, uint8 columns
                   "rtopk::rtopk_wave_kernel<4, 16, 1, true, 1, false, int, 0>",     # M = 4096
                   "rtopk::rtopk_wave_kernel<4, 1, 8, true, 1, false, int, 2>",      # bfloat16 rows, M = 256
                   "rtopk::rtopk_dense_kernel<4, 1, 4, true, 1>",
                   "rtopk::rtopk_wave_kernel<4, 1, 8, true, 1, false, unsigned char, 0>",  # byte-wide columns keep 8 rows
                   "rtopk::rtopk_block_kernel<4, 16, 8, 1, false, 0, false>",        # M = 32768
                   "rtopk::rtopk_stream_kernel<4, 1, false>",                        # M > 65536
                   "rtopk::maxk_scatter_rows_kernel<int, 8, true>",
                   "rtopk::maxk_gather_rows_kernel<unsigned char, 8, true>"):
        assert needle in syms, needle
