"""Host-code sanitizer pass: the offline packer and the C oracle are compiled with
-fsanitize=address,undefined (gcc, CPU only) together with tests/native/sanitize_roundtrip.cpp
and run through a pack / unpack / dequantise / multiply round trip and their error paths."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_01229_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_packer_and_c_oracle_under_asan_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_o = str(tmp_path / "lqq_oracle.o")
    exe = str(tmp_path / "sanitize_roundtrip")
    # the oracle's OpenMP pragmas are left off here: one thread, same arithmetic
    subprocess.run(["gcc", "-std=c11", *san, "-Wno-unknown-pragmas", "-c", os.path.join(ROOT, "oracle", "lqq_oracle.c"),
                    "-o", oracle_o], check=True)
    subprocess.run(["g++", "-std=c++17", *san, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                    os.path.join(ROOT, "tests", "native", "sanitize_roundtrip.cpp"), os.path.join(CSRC, "lqq_pack.cpp"),
                    oracle_o, "-static-libasan", "-static-libubsan", "-lpthread", "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "sanitize_roundtrip ok" in res.stdout
