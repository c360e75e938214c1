"""CPU-only sanitizer target: the oracle, the input generator and the library's host-side shape
classification are compiled with -fsanitize=address,undefined (no recovery) into one program
(tests/sanitize_main.cpp) that replays the Algorithm 2 hand traces, checks the exact-mode functions
against a stable sort on tiny tie-heavy rows, and sweeps the classification over every row width.
Nothing here runs on a GPU, and no GPU code is ever built with a sanitizer."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_generator_and_shape_classification_under_asan_ubsan(tmp_path):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = tmp_path / "sanitize_main"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "paper_2409_00822_amd", "csrc"),
           os.path.join(ROOT, "tests", "sanitize_main.cpp"), os.path.join(ROOT, "oracle", "rtopk_oracle.cpp"),
           os.path.join(ROOT, "workloads", "gen.cpp"), "-o", str(exe)]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "cannot find" in built.stderr and "san" in built.stderr:
        pytest.skip("static sanitizer runtimes are not installed")
    assert built.returncode == 0, built.stderr[-3000:]
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([str(exe), os.path.join(ROOT, "tests", "golden", "alg2_handtrace.txt")], capture_output=True,
                         text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "failures 0" in run.stdout, run.stdout
    # the sweep really covered every width, the traces and the brute-force rows
    words = run.stdout.replace(",", " ").split()
    assert int(words[words.index("traces") + 1]) >= 16
    assert int(words[words.index("shapes") + 1]) > 65536 * 20
