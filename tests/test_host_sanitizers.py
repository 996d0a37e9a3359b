"""The host half of the library (quantiser, index builder, chunk order) compiled with AddressSanitizer and
UndefinedBehaviorSanitizer and driven directly on random shapes.  Host code only; no GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "host_sanitizer")
    cmd = [gxx, "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_1509_05186_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_sanitizer_main.cpp"), os.path.join(ROOT, "paper_1509_05186_amd", "csrc", "etf_host.cpp"),
           "-pthread", "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0 and "sanitize" in res.stdout and ("cannot find" in res.stdout or "unrecognized" in res.stdout):
        pytest.skip("this g++ has no sanitizer runtime")
    assert res.returncode == 0, res.stdout
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert run.returncode == 0 and "host sanitizer run: ok" in run.stdout, run.stdout[-3000:]
