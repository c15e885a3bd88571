"""The library's host side (configuration checks, scratch-layout arithmetic, launch planner,
argument validation) built with AddressSanitizer and UndefinedBehaviorSanitizer and driven
through ordinary, edge and hostile inputs by tests/host/sanitize_driver.cpp.  Host code only:
the device code is compiled as usual and never runs here."""
import os
import shutil
import subprocess

import pytest

from paper_2512_04857_amd import build as libbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which(libbuild.hipcc()) is None, reason="hipcc not found")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    lib = tmp_path / "liblinear_kv_san.so"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    flags = [f for f in libbuild.FLAGS if f != "-O3"] + ["-O1"]
    srcs = [os.path.join(libbuild.CSRC, s) for s in libbuild.SOURCES]
    subprocess.run([libbuild.hipcc(), *flags, *libbuild.PRELOAD, *san, *srcs, "-o", str(lib)], check=True,
                   capture_output=True, timeout=900)
    exe = tmp_path / "sanitize_driver"
    subprocess.run([libbuild.hipcc(), "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
                    "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "host", "sanitize_driver.cpp"), "-L", str(tmp_path),
                    "-llinear_kv_san", f"-Wl,-rpath,{tmp_path}", "-o", str(exe)], check=True, capture_output=True,
                   timeout=300)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600, env=env)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-4000:]
    assert "sanitize_driver ok" in p.stdout
