"""AddressSanitizer + UndefinedBehaviorSanitizer runs of host code (no GPU): the CPU oracle on small inputs with edge
cases, and the library's index-file loader on good and malformed files.  The sanitizers are compiled into host code
only; device code is built as usual and never runs here."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
PKG = os.path.join(ROOT, "paper_2503_14649_amd")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, f"{' '.join(cmd)}\n{p.stdout[-4000:]}"
    return p.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_check")
    _run(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          os.path.join(NATIVE, "oracle_sanitize_check.c"), os.path.join(ROOT, "oracle", "rago_oracle.c"), "-lm", "-o", exe])
    out = _run([exe], env=ENV, timeout=300)
    assert "oracle sanitize check ok" in out


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_index_file_loader_is_clean_under_asan_and_ubsan(tmp_path):
    """The translation unit that holds the loader is rebuilt with host sanitizers and linked in front of the shipped
    library (which supplies the kernels' launchers), so the loader that runs is the instrumented one."""
    lib = os.path.join(PKG, "librago.so")
    if not os.path.exists(lib):
        from paper_2503_14649_amd import build
        build.build()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    common = ["hipcc", "-O1", "-g", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Xclang", "-target-feature",
              "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unused-value", "-I" + os.path.join(ROOT, "include")]
    api_o, drv_o, exe = str(tmp_path / "api_san.o"), str(tmp_path / "drv.o"), str(tmp_path / "loader_sanitize_check")
    _run([*common, *san, "-c", os.path.join(PKG, "csrc", "api.hip"), "-o", api_o])
    _run([*common, *san, "-c", "-x", "hip", os.path.join(NATIVE, "loader_sanitize_check.cpp"), "-o", drv_o])
    _run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", drv_o, api_o,
          "-L" + PKG, "-lrago", "-Wl,-rpath," + PKG, "-o", exe])
    files = tmp_path / "files"
    files.mkdir()
    out = _run([exe, str(files)], env=ENV, timeout=300)
    assert "loader sanitize check ok" in out
