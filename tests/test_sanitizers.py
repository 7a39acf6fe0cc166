"""CPU builds under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU involved):
the C oracle on small shapes, and the host side of the C-ABI library (argument checks, size
arithmetic, dispatch predicates) on calls that are refused before any launch."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)          # the sanitizer runtime has to come first in the process


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
                    os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "bra_oracle.c"),
                    "-o", exe, "-lm"], check=True)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="hipcc not found")
def test_library_host_code_under_sanitizers(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2303_08810_amd import build as bra_build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    objs = bra_build.compile_objects(tag="host_sanitize", extra_flags=["-g"] + host, opt="-O1")
    exe, drv = str(tmp_path / "api_driver"), str(tmp_path / "api_driver.o")
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-c", os.path.join(HERE, "api_driver.cpp"), "-o", drv], check=True)
    subprocess.run([hipcc, "--offload-arch=gfx950", drv] + objs + ["-fsanitize=address,undefined", "-o", exe],
                   check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
