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


def test_binding_fails_loudly_without_the_library(tmp_path):
    """The product path has no fallback: a copy of the package without libraggedshard.so cannot be
    imported, and the message names the build step."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2602_22437_amd"
    pkg.mkdir()
    for name in ("__init__.py", "binding.py"):
        shutil.copy(os.path.join(ROOT, "paper_2602_22437_amd", name), pkg / name)
    r = subprocess.run([sys.executable, "-c", "import paper_2602_22437_amd.binding"], cwd=tmp_path,
                       capture_output=True, text=True, timeout=120,
                       env={k: v for k, v in os.environ.items() if k != "PYTHONPATH"})
    assert r.returncode != 0
    assert "ImportError" in r.stderr and "libraggedshard.so is missing" in r.stderr and "no fallback" in r.stderr


def test_product_code_never_touches_the_oracle():
    """oracle/ is test infrastructure: nothing in the package imports it, and bench.py does so only
    inside its CPU-baseline leg."""
    import re
    pkg = os.path.join(ROOT, "paper_2602_22437_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "oracle/" not in text and "liboracle" not in text, f
    bench = open(os.path.join(ROOT, "bench.py")).read()
    top_level = [l for l in bench.splitlines() if re.match(r"(from|import)\s+oracle\b", l)]
    assert top_level == []          # only function-local imports, in _cpu_sample / cpu_baseline*
    for m in re.finditer(r"^( +)(from|import)\s+oracle\b", bench, re.M):
        before = bench[:m.start()]
        func = re.findall(r"^def (\w+)", before, re.M)[-1]
        assert func in ("_cpu_sample", "cpu_baseline", "cpu_baseline_all_cores"), func
