"""include/raggedshard.h is a C header: tests/c_abi/check.c is compiled as strict C99 against it,
linked with the built library and run on the host half of the interface (no GPU needed)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2602_22437_amd")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_header_compiles_as_c99_and_host_calls_work(tmp_path):
    lib = os.path.join(PKG, "libraggedshard.so")
    assert os.path.exists(lib), "build the library first"
    exe = str(tmp_path / "c_abi_check")
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi", "check.c"), "-L", PKG, "-lraggedshard",
           "-Wl,-rpath," + PKG, "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), (run.stdout[-1000:], run.stderr[-2000:])
