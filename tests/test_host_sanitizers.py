"""The host-only entry points under AddressSanitizer + UndefinedBehaviorSanitizer (a separate build of
plan.cpp, balance.cpp and auto_select.cpp with the C++ driver tests/host_sanitize_main.cpp)."""
import os
import shutil
import subprocess
import tempfile

import pytest

from paper_2503_07680_amd import build as B

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_entry_points_are_clean_under_asan_and_ubsan():
    srcs = [os.path.join(B.CSRC, f) for f in ("plan.cpp", "balance.cpp", "auto_select.cpp")]
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_sanitize")
        cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=all", "-I", B.INCLUDE, os.path.join(HERE, "host_sanitize_main.cpp")] + srcs + ["-o", exe]
        subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        # the link-order check is off because the environment may preload a library of its own
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
        r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, env=env, timeout=300)
        assert r.returncode == 0 and r.stdout.decode().strip().endswith("ok"), r.stdout.decode()[-3000:]
