"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code: the C oracle (all of it) and the host
pass of the library sources (argument validation, workspace carving, launch planning -- everything before the first
kernel launch).  Each build is driven by a small program under tests/sanitize/ whose exit status is the verdict.
No GPU is used: the GPU code objects are compiled without sanitizers and never run here."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
# the container preloads a small library of its own ahead of the sanitizer runtime; that order is harmless
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe):
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, f"{exe} failed ({r.returncode}):\n{r.stdout}\n{r.stderr}"
    return r.stdout


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-o", exe,
                    os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "st_oracle.c"), "-lm"], check=True)
    assert "ok" in _run(exe)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_library_host_code_under_address_and_ub_sanitizers(tmp_path):
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
             "-fno-sanitize-recover=all", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    csrc = os.path.join(ROOT, "paper_2504_12329_amd", "csrc")
    from paper_2504_12329_amd import build as lib_build
    srcs = [os.path.join(csrc, f) for f in lib_build.SOURCES]
    srcs.append(os.path.join(SAN, "abi_driver.cpp"))

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run(["hipcc", *flags, "-x", "hip", "-c", src, "-o", obj], check=True, capture_output=True)
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, srcs))
    exe = str(tmp_path / "abi_san")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", exe, *objs],
                   check=True, capture_output=True)
    assert "ok" in _run(exe)
