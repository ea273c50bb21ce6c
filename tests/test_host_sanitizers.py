"""The host half of libkvswitch (plain C++) under AddressSanitizer and UndefinedBehaviorSanitizer:
tests/host_sanitize_driver.cpp is compiled with the two host sources and run.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2403_11805_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"),
           os.path.join(CSRC, "kv_host.cpp"), os.path.join(CSRC, "kv_lctru.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    # the environment is inherited as it is; ASan is told not to insist on being the first library
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "host sanitizer drive ok" in res.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_from_several_threads_under_tsan(tmp_path):
    """Six threads call the pure host functions at once and each drives a queue of its own:
    ThreadSanitizer reports no race, every thread sees its own error text."""
    exe = str(tmp_path / "host_threads")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=thread", "-pthread",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_threads_driver.cpp"),
           os.path.join(CSRC, "kv_host.cpp"), os.path.join(CSRC, "kv_lctru.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1:exitcode=66")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    if "FATAL: ThreadSanitizer" in res.stderr and "unexpected memory mapping" in res.stderr:
        pytest.skip("ThreadSanitizer cannot map its shadow memory in this container")
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "host threads drive ok" in res.stdout
