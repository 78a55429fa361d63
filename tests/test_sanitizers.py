"""Host code under AddressSanitizer + UBSan: the CPU oracle and the library's host-only segment-table
code are compiled with gcc's sanitizers into a small driver (tests/sanitize_host.cpp) and run on ragged
inputs.  No GPU code is involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_oracle_and_segment_table_are_clean_under_asan_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-O1", "-g"]
    obj = str(tmp_path / "oracle.o")
    exe = str(tmp_path / "sanitize_host")
    subprocess.run(["gcc", "-std=c99", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "adagc_oracle.c"),
                    "-o", obj] + san, check=True)
    subprocess.run(["g++", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "sanitize_host.cpp"),
                    os.path.join(ROOT, "paper_2502_11034_amd", "csrc", "segment_table.cpp"), obj, "-o", exe, "-lm"] + san,
                   check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)       # the sanitizer runtime must come first
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "sanitize_host: ok" in res.stdout
