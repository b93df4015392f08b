"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU side: the oracle, and the host-only
paths of libtidal (configuration, arena layout, copy plan, LoRA launch plan, argument validation,
state machine) built from the library's own sources with the kernel launchers replaced by stand-ins.

Both are small C / C++ programs under tests/sanitize/ that run everything on seeded inputs and check
their invariants with plain ifs; the sanitizers turn any out-of-bounds access, use after free or
undefined operation into a non-zero exit status.  No GPU is involved (device code is compiled but
never runs; GPU sanitizers are not used).
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
CSRC = os.path.join(ROOT, "paper_2503_06421_amd", "csrc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, **kw)


def check_clean(p, marker):
    out = p.stdout + p.stderr
    assert p.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert marker in p.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    p = run(["gcc", "-std=c99", "-O1", "-g", "-mfma", "-ffp-contract=off", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-o", exe,
             os.path.join(ROOT, "oracle", "tidal_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-lm"])
    assert p.returncode == 0, p.stderr[-4000:]
    check_clean(run([exe], env=ENV), "oracle sanitizer run ok")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_host_paths_of_libtidal_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"):
        host_san += ["-Xarch_host", f]                       # host code only: GPU sanitizers are not available here
    p = run(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san,
             "-I", os.path.join(ROOT, "include"), "-I", CSRC,
             os.path.join(CSRC, "tidal.cpp"), os.path.join(CSRC, "tidal_lora.cpp"), os.path.join(CSRC, "tidal_apply.cpp"),
             os.path.join(CSRC, "plan.cpp"),
             os.path.join(SAN, "launch_stubs.cpp"), os.path.join(SAN, "host_driver.cpp"),
             "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-pthread", "-o", exe])
    assert p.returncode == 0, p.stderr[-4000:]
    check_clean(run([exe], env=ENV), "host sanitizer run ok")
