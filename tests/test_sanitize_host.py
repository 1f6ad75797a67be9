"""AddressSanitizer / UndefinedBehaviorSanitizer runs of the CPU-side code: the host-only translation unit
of the C ABI's argument validation and workspace carving, and the fp64 oracle.  (GPU code cannot run under
a sanitizer here; these are the parts of the build that run on the host.)"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
# (the link-order check is off: a preloaded library in the environment would otherwise stop the program at start)
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")


def _build_and_run(tmp_path, compiler, sources, extra):
    if shutil.which(compiler) is None:
        pytest.skip(compiler + " not available")
    exe = str(tmp_path / "check")
    cmd = [compiler] + SAN + extra + sources + ["-o", exe, "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    run = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert run.returncode == 0, (run.stdout[-1000:], run.stderr[-3000:])
    assert run.stdout.startswith("ok"), run.stdout
    return run.stdout


def test_abi_validation_and_workspace_carving_under_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "g++", [os.path.join(ROOT, "tests", "sanitize", "host_layout_check.cc")],
                         ["-std=c++17", "-I", os.path.join(ROOT, "include"),
                          "-I", os.path.join(ROOT, "paper_2506_16640_amd", "csrc")])
    assert int(out.split()[1]) > 10000


def test_oracle_under_sanitizers(tmp_path):
    _build_and_run(tmp_path, "gcc", [os.path.join(ROOT, "tests", "sanitize", "oracle_check.c"),
                                     os.path.join(ROOT, "oracle", "entmax_oracle.c")], ["-std=c11", "-fopenmp"])
