"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (host pass only;
the device code is compiled as always and no GPU is touched): a C++ driver runs the scheduling
round on random prefix-sharing streams with store / evict events, the threshold routines and the
argument checks of every GPU entry point against a sanitized build of the library."""
import os
import shutil
import subprocess
import tempfile

import pytest

from paper_2605_02960_amd import build as moe_build

HERE = os.path.dirname(os.path.abspath(__file__))
SAN = ("-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined", "-g")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_host_code_is_clean_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory(prefix="moe_san_") as tmp:
        lib = moe_build.build(extra=SAN, out=os.path.join(tmp, "libmoeprefill_san.so"), link_extra=SAN)
        exe = os.path.join(tmp, "sanitize_driver")
        subprocess.check_call(["hipcc", "-O1", "-g", "-std=c++17", "-x", "c++", "-fsanitize=address",
                               "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                               os.path.join(HERE, "host", "sanitize_driver.cpp"), "-x", "none", lib,
                               "-Wl,-rpath," + tmp, "-o", exe])
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
        assert p.returncode == 0, p.stdout[-4000:]
        assert "sanitize_driver: ok" in p.stdout and "ERROR: AddressSanitizer" not in p.stdout \
            and "runtime error" not in p.stdout, p.stdout[-4000:]
