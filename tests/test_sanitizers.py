"""Host code under AddressSanitizer and UBSan (CPU only): the oracle and the
schedule builder, compiled with gcc/g++ -fsanitize=address,undefined together
with small drivers that walk every table and compare against the definition."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def build_and_run(tmp_path, compiler, std, sources, name):
    exe = str(tmp_path / name)
    res = subprocess.run([compiler, std, *SAN, "-I", os.path.join(ROOT, "include"), *sources, "-o", exe],
                         capture_output=True, text=True)
    if res.returncode != 0 and "sanitize" in res.stderr:
        pytest.skip("sanitizer runtime not available: " + res.stderr[-200:])
    assert res.returncode == 0, res.stderr
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    return out.stdout


def test_oracle_is_clean_under_asan_ubsan(tmp_path):
    out = build_and_run(tmp_path, "gcc", "-std=c11",
                        [os.path.join(ROOT, "tests", "c", "oracle_sanitize.c"),
                         os.path.join(ROOT, "oracle", "sparbit_oracle.c")], "oracle_sanitize")
    assert "bad=0" in out


def test_schedule_builder_is_clean_under_asan_ubsan(tmp_path):
    out = build_and_run(tmp_path, "g++", "-std=c++17",
                        [os.path.join(ROOT, "tests", "c", "plan_sanitize.cpp"),
                         os.path.join(ROOT, "paper_2109_08751_amd", "csrc", "plan.cpp")], "plan_sanitize")
    assert out.startswith("ok")
