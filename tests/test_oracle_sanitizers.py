"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small C++ driver
(tests/oracle_sanitizer_drive.cpp) includes oracle/bct_ref.cpp, calls every entry point on exact-size heap
buffers (both dtypes, GQA, shared and per-sequence keys, read-only / write-only / gated steps and chunks,
export / import, per-sequence swap) and must finish without a report."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "drive")
    cc = ["g++", "-std=c++17", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", os.path.join(HERE, "oracle_sanitizer_drive.cpp"),
          "-o", exe]
    r = subprocess.run(cc, capture_output=True, text=True)
    if r.returncode != 0 and "cannot find" in r.stderr and "asan" in r.stderr:
        pytest.skip("the sanitizer runtimes are not installed")
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    if r.returncode != 0 and "ASan runtime does not come first" in r.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from loading first")
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "oracle sanitizer drive: ok" in r.stdout
