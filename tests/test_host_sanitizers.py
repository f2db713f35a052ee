"""The host-side Reuse Store under AddressSanitizer, UBSan and ThreadSanitizer
(CPU only): tests/host_fuzz.cpp drives random histories with every plan flag."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ is not installed")
def test_random_histories_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", os.path.join(HERE, "host_fuzz.cpp"),
           os.path.join(ROOT, "paper_2512_01357_amd", "csrc", "reuse_store.cpp"), "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    out = subprocess.run([exe, "24"], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         timeout=300)
    assert out.returncode == 0, out.stdout[-4000:]
    assert "ok 24 histories" in out.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ is not installed")
def test_stores_on_several_threads_share_nothing_under_tsan(tmp_path):
    exe = str(tmp_path / "host_fuzz_tsan")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-fno-omit-frame-pointer", "-pthread",
           os.path.join(HERE, "host_fuzz.cpp"),
           os.path.join(ROOT, "paper_2512_01357_amd", "csrc", "reuse_store.cpp"), "-o", exe]
    subprocess.check_call(cmd)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)
    env["TSAN_OPTIONS"] = "halt_on_error=1"
    out = subprocess.run([exe, "16", "4"], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         timeout=300)
    assert out.returncode == 0, out.stdout[-4000:]
    assert "ok 16 histories" in out.stdout
