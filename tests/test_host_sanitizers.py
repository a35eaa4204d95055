"""Host code of the library (the compressor) and the oracle under AddressSanitizer and
UndefinedBehaviorSanitizer: a small C++ driver is compiled with g++ together with
endor_host.cpp and endor_oracle.c and run on ragged shapes with exactly sized buffers."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_compressor_and_oracle_under_asan_ubsan(tmp_path):
    exe = tmp_path / "host_sanitizer_driver"
    obj = tmp_path / "oracle.o"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
                           "-c", os.path.join(ROOT, "oracle", "endor_oracle.c"), "-o", str(obj)])
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-pthread", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2406_11674_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
                           os.path.join(ROOT, "paper_2406_11674_amd", "csrc", "endor_host.cpp"),
                           str(obj), "-o", str(exe)])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    proc = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert proc.returncode == 0, proc.stdout
    assert proc.stdout.strip().startswith("ok"), proc.stdout
