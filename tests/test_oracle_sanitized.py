"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): oracle/sanitize_check.cpp
drives every oracle function over the hand-computed case and ragged random shapes; any report fails the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-o", exe, os.path.join(ROOT, "oracle", "sanitize_check.cpp")])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "sanitize_check ok" in r.stdout, r.stdout + r.stderr
