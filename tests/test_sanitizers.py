"""Host code and oracle under AddressSanitizer + UndefinedBehaviorSanitizer.

Builds the host-only translation unit of libkvm (free list, divider, validation,
helpers) and the C oracle with -fsanitize=address,undefined and runs seeded random
drivers over them (tests/sanitize/).  GPU sanitizers are not available on the
target boxes; the kernels' bounds rest on the host-side validation exercised here
and on the in-kernel clamps."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
# the environment is passed on as it is; a preloaded library ahead of the sanitizer
# runtime is tolerated instead of being removed
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="halt_on_error=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, **kw)
    assert r.returncode == 0, "%s\n%s" % (" ".join(cmd), r.stdout[-4000:])
    return r.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_host_code_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_driver")
    run(["g++", "-std=c++17"] + SAN + ["-I" + os.path.join(ROOT, "include"),
                                        "-I" + os.path.join(ROOT, "paper_2501_06709_amd", "csrc"),
                                        os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
                                        os.path.join(ROOT, "paper_2501_06709_amd", "csrc", "kvm_host.cpp"),
                                        "-o", exe])
    assert "host driver ok" in run([exe], env=ENV)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host compiler")
def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    run(["gcc", "-std=c99"] + SAN + [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                                     os.path.join(ROOT, "oracle", "kvm_oracle.c"), "-o", exe, "-lm"])
    assert "oracle driver ok" in run([exe], env=ENV)
