"""Multiply-high division of the GPU library's row bookkeeping, built for the host (CPU only): the quotient
must equal plain integer division for every dividend below 2^31 the checker tries (all small divisors, divisors
around powers of two, random large ones; dividends around multiples of the divisor and at the top of the range)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def test_fast_division_matches_plain_division(tmp_path):
    exe = str(tmp_path / "fastdiv_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-o", exe, os.path.join(HERE, "fastdiv_check.cpp")], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout + r.stderr
