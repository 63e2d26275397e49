"""The host half of the library (offline quantization, packing, unpacking, adapters: csrc/prepare.cpp) built with the
host compiler under AddressSanitizer + UndefinedBehaviorSanitizer and driven over small ragged shapes, with every output
buffer sized exactly as the *_prepared_sizes calls report.  No GPU code takes part."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.timeout(600)
def test_prepare_pack_unpack_under_asan_and_ubsan(tmp_path):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path / "host_sanitize")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "paper_2411_05007_amd", "csrc", "prepare.cpp"), os.path.join(HERE, "host_sanitize_driver.cpp"),
           "-o", exe, "-lpthread"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    # a preloaded library ahead of the sanitizer runtime is fine here; leaks are errors, as is any report
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    run = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=500)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "all ok" in run.stdout
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr
