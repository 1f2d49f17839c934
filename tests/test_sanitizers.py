"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU, no device code sanitised).

The oracle: a small C++ driver (tests/oracle_sanitizer_drive.cpp) includes oracle/bct_ref.cpp, calls every
entry point on exact-size heap buffers (both dtypes, GQA, shared and per-sequence keys, read-only /
write-only / gated steps and chunks, export / import, per-sequence swap) and must finish without a report.

The library's host layer: csrc/*.hip compiled with the sanitizers on the host pass only and linked with
tests/host_sanitizer_drive.cpp, which walks the size queries, the launch planning and the argument checks
that return before any GPU call."""
import concurrent.futures
import glob
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


HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_library_host_layer_is_clean_under_asan_and_ubsan(tmp_path):
    root = os.path.dirname(HERE)
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I", os.path.join(root, "include")]
    # host pass only: every sanitizer option directly after -Xarch_host
    flags += "-Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined".split()
    srcs = sorted(glob.glob(os.path.join(root, "paper_2411_15785_amd", "csrc", "*.hip")))
    assert srcs

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        extra = ["-x", "hip"] if src.endswith(".cpp") else []
        r = subprocess.run([HIPCC, *flags, *extra, "-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return obj

    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, srcs + [os.path.join(HERE, "host_sanitizer_drive.cpp")]))
    exe = str(tmp_path / "host_drive")
    link = "-fsanitize=address -fsanitize=undefined -fno-gpu-sanitize".split()   # host runtimes only
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-rdc", *link, *objs, "-o", exe],
                       capture_output=True, text=True)
    if r.returncode != 0 and "asan" in r.stderr and "cannot find" in r.stderr:
        pytest.skip("the sanitizer runtimes are not installed")
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    if r.returncode != 0 and "ASan runtime does not come first" in r.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from loading first")
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "host sanitizer drive: ok" in r.stdout
