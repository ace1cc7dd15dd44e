"""Native CPU checks of host code, built with plain g++ (no GPU toolchain, nothing launched):
  * tests/cpp/sanitize_host.cpp links csrc/host_ops.cpp and oracle/kvbfp_oracle.cpp into one program
    under AddressSanitizer + UndefinedBehaviorSanitizer and walks every host entry point and oracle
    function, edge cases and error paths included;
  * tests/cpp/fastdiv_check.cpp checks the multiply-shift division of the cache-write kernel
    (csrc/fastdiv.h) against plain division over the whole numerator range it is used for."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2403_20137_amd", "csrc")]

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")


def _build_and_run(tmp_path, name, sources, flags, timeout):
    exe = str(tmp_path / name)
    cmd = ["g++", "-std=c++17", *flags, *INC, *[os.path.join(ROOT, s) for s in sources], "-o", exe]
    subprocess.run(cmd, check=True, timeout=300)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=timeout, env=env)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    return r.stdout


def test_host_code_and_oracle_under_address_and_ub_sanitizers(tmp_path):
    out = _build_and_run(
        tmp_path, "sanitize_host",
        ["tests/cpp/sanitize_host.cpp", "paper_2403_20137_amd/csrc/host_ops.cpp", "oracle/kvbfp_oracle.cpp"],
        ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
         "-frounding-math"], timeout=120)
    assert "sanitize_host ok" in out


def test_fastdiv_is_exact_below_two_to_the_31(tmp_path):
    out = _build_and_run(tmp_path, "fastdiv_check", ["tests/cpp/fastdiv_check.cpp"], ["-O2"], timeout=300)
    assert "fastdiv ok" in out
