"""The C ABI driven from a plain C program (tests/abi_errors.c): every error path returns its code, nothing crashes."""
import os
import subprocess

import pytest

from paper_2412_04788_amd import guide

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build(tmp_path):
    exe = tmp_path / "abi_errors"
    lib_dir = os.path.dirname(guide.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "abi_errors.c"), "-o", str(exe),
                           "-L", lib_dir, "-l:libguide.so", "-Wl,-rpath," + lib_dir])
    return str(exe)


def test_error_paths_without_a_context(tmp_path):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: the full program runs in the gpu test")
    r = subprocess.run([_build(tmp_path), "nogpu"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "0 failure(s)" in r.stdout and r.stdout.count("ok ") >= 17


@pytest.mark.gpu
def test_error_paths_on_the_gpu(tmp_path):
    r = subprocess.run([_build(tmp_path)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "0 failure(s)" in r.stdout and r.stdout.count("ok ") >= 60
